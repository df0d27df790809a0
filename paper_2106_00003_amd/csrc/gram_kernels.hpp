// Gram matrix of the reverse sweep for wide batches: C = Y G^T (rows x rows, contraction over the B columns).
//
// Why it is on the path.  The reverse sweep's per-pair sums (paper Section 4.1/4.2: the row sums of the matrix A,
// the only step of the method that reduces across data) are entries of z gbar^T = A_k (Y G^T) A_k^T, where A_k is
// the product of the transposed blocks undone so far.  For B >= 2n it is cheaper to contract over B once, here,
// and to run the sweep on the rows x rows operand C instead of on all B columns.  This is the one dense
// contraction of the library, so it runs on the matrix cores: float32 MFMA (v_mfma_f32_32x32x2_f32), float32
// accumulation, no reduced-precision inputs.
//
// Kernel.  Both operands are row-major rows x B, i.e. contiguous along the contraction index.  A workgroup of
// four wavefronts computes a 128 x 128 tile of C for one slice of the contraction range; each wavefront owns a
// 64 x 64 quarter as 2 x 2 MFMA tiles of 32 x 32 (64 accumulator registers).  Per step of kGramK = 32 columns the
// workgroup brings a 128 x 32 panel of Y and of G from memory into LDS (16-byte loads, staged through registers
// one step ahead, two LDS buffers), and every lane reads its MFMA operands from LDS as 16-byte vectors: lane l
// takes row l % 32 of the panel and the four columns 4 * (l / 32) + 8 j .. + 3 for j = 0..3, so that the s-th
// of the 16 MFMAs of a step (K = 2 each) contracts columns {8 j + s', 8 j + 4 + s'} (j = s / 4, s' = s % 4) --
// a permutation of the step's 32 columns that is the same for both operands.  Rows of a panel are padded to 36
// floats in LDS so that the 16-byte accesses of a quarter wavefront fall in distinct banks.
// The contraction range is cut into `slices` (split-K): slice s writes its own rows x rows matrix and
// sum_slices_kernel adds them in slice order, so the result does not depend on scheduling.
#pragma once
#include <hip/hip_runtime.h>

namespace givens {

constexpr int kGramTile = 128;   // tile of C per workgroup
constexpr int kGramK = 32;       // contraction columns per step
constexpr int kGramPitch = 36;   // floats per panel row in LDS
constexpr int kGramThreads = 256;

typedef float gram_acc_t __attribute__((ext_vector_type(16)));

struct GramPanels {
    float y[2][kGramTile * kGramPitch];
    float g[2][kGramTile * kGramPitch];
};

// One thread's share of a 128 x 32 panel: four 16-byte pieces; piece i is row (t + 256 i) / 8, columns
// 4 * ((t + 256 i) % 8) .. + 3.  Rows beyond `rows` and columns beyond `kend` read as zero.
__device__ __forceinline__ void gram_fetch(float4 (&dst)[4], const float *__restrict__ src, long long ld, int rows,
                                           int row0, long long k0, long long kend, int vec_ok)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = (int)threadIdx.x + kGramThreads * i;
        const int r = row0 + (c >> 3);
        const long long k = k0 + 4 * (c & 7);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < rows) {
            const float *p = src + (long long)r * ld + k;
            if (vec_ok && k + 4 <= kend) {
                v = *reinterpret_cast<const float4 *>(p);
            } else {
                if (k < kend) v.x = p[0];
                if (k + 1 < kend) v.y = p[1];
                if (k + 2 < kend) v.z = p[2];
                if (k + 3 < kend) v.w = p[3];
            }
        }
        dst[i] = v;
    }
}
__device__ __forceinline__ void gram_stash(float *panel, const float4 (&src)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = (int)threadIdx.x + kGramThreads * i;
        *reinterpret_cast<float4 *>(panel + (c >> 3) * kGramPitch + 4 * (c & 7)) = src[i];
    }
}

// C_s[i][j] = sum over the slice's columns b of Y[i][b] * G[j][b]; grid = (tiles, tiles, slices).
// C has room for gridDim.z matrices of rows x rows floats.
__global__ __launch_bounds__(kGramThreads, 2) void gram_tile_kernel(int rows, long long B, long long slice_cols,
                                                                    const float *__restrict__ Y,
                                                                    const float *__restrict__ G, float *__restrict__ C,
                                                                    int vec_ok)
{
    __shared__ GramPanels sh;
    const int tile_i = blockIdx.y, tile_j = blockIdx.x;
    const long long kbeg = (long long)blockIdx.z * slice_cols;
    const long long kend = (kbeg + slice_cols < B) ? kbeg + slice_cols : B;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = (wave >> 1) * 64, wj = (wave & 1) * 64;        // this wavefront's quarter of the tile
    const int frag_row = lane & 31, frag_col = 4 * (lane >> 5);

    gram_acc_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    float4 ry[4], rg[4];
    gram_fetch(ry, Y, B, rows, tile_i * kGramTile, kbeg, kend, vec_ok);
    gram_fetch(rg, G, B, rows, tile_j * kGramTile, kbeg, kend, vec_ok);
    int buf = 0;
    for (long long k0 = kbeg; k0 < kend; k0 += kGramK, buf ^= 1) {
        gram_stash(sh.y[buf], ry);
        gram_stash(sh.g[buf], rg);
        __syncthreads();   // this step's panels are in LDS; the other buffer is free (its readers passed this barrier)
        if (k0 + kGramK < kend) {
            gram_fetch(ry, Y, B, rows, tile_i * kGramTile, k0 + kGramK, kend, vec_ok);
            gram_fetch(rg, G, B, rows, tile_j * kGramTile, k0 + kGramK, kend, vec_ok);
        }
        const float *py = sh.y[buf] + (wi + frag_row) * kGramPitch + frag_col;
        const float *pg = sh.g[buf] + (wj + frag_row) * kGramPitch + frag_col;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 y0 = *reinterpret_cast<const float4 *>(py + 8 * j);
            const float4 y1 = *reinterpret_cast<const float4 *>(py + 32 * kGramPitch + 8 * j);
            const float4 g0 = *reinterpret_cast<const float4 *>(pg + 8 * j);
            const float4 g1 = *reinterpret_cast<const float4 *>(pg + 32 * kGramPitch + 8 * j);
            const float ya[2][4] = {{y0.x, y0.y, y0.z, y0.w}, {y1.x, y1.y, y1.z, y1.w}};
            const float ga[2][4] = {{g0.x, g0.y, g0.z, g0.w}, {g1.x, g1.y, g1.z, g1.w}};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(ya[a][s], ga[b][s], acc[a][b], 0, 0, 0);
        }
    }

    // accumulator layout of the 32 x 32 MFMA: register v of lane l is row 8 (v / 4) + 4 (l / 32) + v % 4,
    // column l % 32 of the tile
    float *out = C + (long long)blockIdx.z * rows * rows;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = tile_j * kGramTile + wj + 32 * b + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = tile_i * kGramTile + wi + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < rows && col < rows) out[(long long)row * rows + col] = acc[a][b][v];
            }
        }
}

// c[0] += c[1] + ... + c[slices-1] element by element, in that order
__global__ void sum_slices_kernel(long long count, int slices, float *__restrict__ c)
{
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (long long)gridDim.x * blockDim.x) {
        float acc = c[i];
        for (int s = 1; s < slices; ++s) acc += c[(long long)s * count + i];
        c[i] = acc;
    }
}

// How many slices the contraction is cut into: enough workgroups to give every compute unit a few, and at
// least a few hundred columns per slice.
inline int gram_slices(int rows, long long B, int compute_units)
{
    const long long tiles = (long long)((rows + kGramTile - 1) / kGramTile) * ((rows + kGramTile - 1) / kGramTile);
    long long s = (4LL * compute_units + tiles - 1) / tiles;
    s = s < 16 ? s : 16;
    const long long by_cols = B / 512 > 1 ? B / 512 : 1;
    s = s < by_cols ? s : by_cols;
    return (int)(s > 1 ? s : 1);
}

// Launches C = Y G^T; C must hold slices * rows * rows floats; the result ends in the first rows * rows.
inline void gram_matrix(int rows, long long B, int slices, const float *Y, const float *G, float *C,
                        hipStream_t stream)
{
    const int tiles = (rows + kGramTile - 1) / kGramTile;
    long long slice_cols = (B + slices - 1) / slices;
    slice_cols = (slice_cols + kGramK - 1) / kGramK * kGramK;      // slices start on a step boundary (16-byte loads)
    const int vec_ok = (B % 4 == 0) && (reinterpret_cast<uintptr_t>(Y) % 16 == 0) &&
                       (reinterpret_cast<uintptr_t>(G) % 16 == 0);
    hipLaunchKernelGGL(gram_tile_kernel, dim3(tiles, tiles, slices), dim3(kGramThreads), 0, stream, rows, B, slice_cols,
                       Y, G, C, vec_ok);
    if (slices > 1)
        hipLaunchKernelGGL(sum_slices_kernel, dim3(1024), dim3(256), 0, stream, (long long)rows * rows, slices, C);
}

} // namespace givens
