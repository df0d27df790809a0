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
// 64 x 64 quarter as 2 x 2 MFMA tiles of 32 x 32 (64 accumulator registers).  Per step of kGramK = 16 columns the
// workgroup brings a 128 x 16 panel of Y and of G from memory into LDS (16-byte loads, staged through registers
// one step ahead, two LDS buffers), and every lane reads its MFMA operands from LDS as 16-byte vectors: lane l
// takes row l % 32 of the panel and the four columns 4 * (l / 32) + 8 j .. + 3 for j = 0, 1, so that the s-th
// of the 8 MFMAs of a step (K = 2 each) contracts columns {8 j + s', 8 j + 4 + s'} (j = s / 4, s' = s % 4) --
// a permutation of the step's 16 columns that is the same for both operands.  Rows of a panel are padded by
// four floats in LDS: the operand reads are then free of bank conflicts; the 16-byte stores of the staging step
// still collide a little (a third of the LDS cycles carry a conflict), hidden behind the MFMA pipe, which is busy
// 93 % of the time.  An unpadded layout with the pieces of a row exchanged by two bits of the row number removes
// those conflicts and measures 5 % slower (4.48 against 4.25 ms), so the padding stays.  41 KB of LDS and under 168 registers: three workgroups per
// compute unit, so that one workgroup's staging and barrier hide behind the others' MFMAs (measured: steps of
// 32 columns with two workgroups per compute unit 4.77 ms, this 4.5 ms at rows = 2048, B = 65536).
// The contraction range is cut into `slices` (split-K): slice s writes its own rows x rows matrix and
// sum_slices_kernel adds them in slice order, so the result does not depend on scheduling.
#pragma once
#include <hip/hip_runtime.h>

namespace givens {

constexpr int kGramTile = 128;   // tile of C per workgroup
constexpr int kGramK = 16;       // contraction columns per step
constexpr int kGramPitch = kGramK + 4; // floats per panel row in LDS
constexpr int kGramPieces = kGramK / 8;  // 16-byte pieces of a panel per thread
constexpr int kGramRowPieces = kGramK / 4; // 16-byte pieces per panel row
constexpr int kGramThreads = 256;

typedef float gram_acc_t __attribute__((ext_vector_type(16)));
typedef float gram_vec4 __attribute__((ext_vector_type(4)));   // a 16-byte piece of a panel

struct GramPanels {
    float y[2][kGramTile * kGramPitch];
    float g[2][kGramTile * kGramPitch];
};

// One thread's share of a 128 x 32 panel: four 16-byte pieces; piece i is row (t + 256 i) / 8, columns
// 4 * ((t + 256 i) % 8) .. + 3.  GUARD: rows beyond `rows` and columns beyond `kend` read as zero and unaligned
// operands are read element by element; without it every piece is one unconditional 16-byte load (the launch
// has checked that the tiles and the slices are full and the rows 16-byte aligned).
template <bool GUARD>
__device__ __forceinline__ void gram_fetch(gram_vec4 (&dst)[kGramPieces], const float *__restrict__ src, long long ld, int rows,
                                           int row0, long long k0, long long kend, int vec_ok)
{
#pragma unroll
    for (int i = 0; i < kGramPieces; ++i) {
        const int c = (int)threadIdx.x + kGramThreads * i;
        const int r = row0 + c / kGramRowPieces;
        const long long k = k0 + 4 * (c % kGramRowPieces);
        const float *p = src + (long long)r * ld + k;
        if constexpr (!GUARD) {
            // past the end of the slice (the prefetch runs one step ahead) the last step of the operand is read
            // instead; what it brings is never used
            const long long ks = k0 < kend ? k0 : kend - kGramK;
            dst[i] = *reinterpret_cast<const gram_vec4 *>(src + (long long)r * ld + ks + 4 * (c % kGramRowPieces));
        } else {
            gram_vec4 v = {0.f, 0.f, 0.f, 0.f};
            if (r < rows) {
                if (vec_ok && k + 4 <= kend) {
                    v = *reinterpret_cast<const gram_vec4 *>(p);
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
}
__device__ __forceinline__ void gram_stash(float *panel, const gram_vec4 (&src)[kGramPieces])
{
#pragma unroll
    for (int i = 0; i < kGramPieces; ++i) {
        const int c = (int)threadIdx.x + kGramThreads * i;
        *reinterpret_cast<gram_vec4 *>(panel + (c / kGramRowPieces) * kGramPitch + 4 * (c % kGramRowPieces)) = src[i];
    }
}

// C_s[i][j] = sum over the slice's columns b of Y[i][b] * G[j][b]; grid = (tiles, tiles, slices).
// C has room for gridDim.z matrices of rows x rows floats.
template <bool GUARD>
__global__ __launch_bounds__(kGramThreads, 3) void gram_tile_kernel(int rows, long long B, long long slice_cols,
                                                                    const float *__restrict__ Y,
                                                                    const float *__restrict__ G, float *__restrict__ C,
                                                                    int vec_ok)
{
    __shared__ GramPanels sh;
    // Workgroups are handed to the eight XCDs (each with an L2 of its own) in turn, in launch order.  The tile a
    // workgroup takes is therefore not the one its launch index names: the list of (slice, tile row, tile column)
    // is cut into eight consecutive parts and workgroup L takes entry L / 8 of part L % 8, so that the workgroups
    // that share an L2 at any time work on a few neighbouring tile rows of one slice and reuse each other's panels.
    const unsigned tiles = gridDim.x, total = gridDim.x * gridDim.y * gridDim.z;
    unsigned id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    if (total % 8 == 0) id = (id % 8) * (total / 8) + id / 8;
    const int tile_j = id % tiles, tile_i = (id / tiles) % tiles;
    const unsigned slice = id / (tiles * tiles);
    const long long kbeg = (long long)slice * slice_cols;
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

    // one step of the contraction on the panels in LDS buffer `buf`
    auto contract = [&](int buf) {
        const float *py = sh.y[buf] + (wi + frag_row) * kGramPitch + frag_col;
        const float *pg = sh.g[buf] + (wj + frag_row) * kGramPitch + frag_col;
#pragma unroll
        for (int j = 0; j < kGramK / 8; ++j) {
            const gram_vec4 ya[2] = {*reinterpret_cast<const gram_vec4 *>(py + 8 * j),
                                     *reinterpret_cast<const gram_vec4 *>(py + 32 * kGramPitch + 8 * j)};
            const gram_vec4 ga[2] = {*reinterpret_cast<const gram_vec4 *>(pg + 8 * j),
                                     *reinterpret_cast<const gram_vec4 *>(pg + 32 * kGramPitch + 8 * j)};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(ya[a][s], ga[b][s], acc[a][b], 0, 0, 0);
        }
    };

    // Panels are fetched one step ahead into registers (two steps ahead measured 2 % faster for 100 more
    // registers, which costs the third workgroup per compute unit) and staged into the LDS buffer of their step's parity right before the barrier that opens the step.
    gram_vec4 ry[kGramPieces], rg[kGramPieces];
    gram_fetch<GUARD>(ry, Y, B, rows, tile_i * kGramTile, kbeg, kend, vec_ok);
    gram_fetch<GUARD>(rg, G, B, rows, tile_j * kGramTile, kbeg, kend, vec_ok);
    int buf = 0;
    for (long long k0 = kbeg; k0 < kend; k0 += kGramK, buf ^= 1) {
        gram_stash(sh.y[buf], ry);
        gram_stash(sh.g[buf], rg);
        __syncthreads();   // this step's panels are in LDS; the other buffer is free (its readers passed this barrier)
        gram_fetch<GUARD>(ry, Y, B, rows, tile_i * kGramTile, k0 + kGramK, kend, vec_ok);
        gram_fetch<GUARD>(rg, G, B, rows, tile_j * kGramTile, k0 + kGramK, kend, vec_ok);
        contract(buf);
    }

    // accumulator layout of the 32 x 32 MFMA: register v of lane l is row 8 (v / 4) + 4 (l / 32) + v % 4,
    // column l % 32 of the tile
    float *out = C + (long long)slice * rows * rows;
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
    // full tiles, full steps in every slice, aligned rows: the kernel without bounds checks in its loads
    const bool full = vec_ok && rows % kGramTile == 0 && B % kGramK == 0;
    if (full)
        hipLaunchKernelGGL(gram_tile_kernel<false>, dim3(tiles, tiles, slices), dim3(kGramThreads), 0, stream, rows, B,
                           slice_cols, Y, G, C, vec_ok);
    else
        hipLaunchKernelGGL(gram_tile_kernel<true>, dim3(tiles, tiles, slices), dim3(kGramThreads), 0, stream, rows, B,
                           slice_cols, Y, G, C, vec_ok);
    if (slices > 1)
        hipLaunchKernelGGL(sum_slices_kernel, dim3(1024), dim3(256), 0, stream, (long long)rows * rows, slices, C);
}

} // namespace givens
