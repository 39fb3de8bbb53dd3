// One-time preparation of a weight matrix: its column-major copy.  The matrix-core path checks uncertain ranks
// against exact fp32 logits of single vocabulary columns; in the row-major matrix a column is one element per
// 128-byte line (64 KB of traffic for a column of 512 elements), in the copy it is K adjacent elements.
#include "device_utils.hpp"
#include "launch.hpp"

namespace slimspec {

// Block (vocabulary tile of 64 columns, contraction tile of 64 rows): read rows of M as 128-byte lines, write
// columns of the copy as 128-byte lines; the tile turns in shared memory (rows padded by one element pair).
__global__ __launch_bounds__(256) void transpose_weights_kernel(
    const uint16_t *__restrict__ M, int K, int V, uint16_t *__restrict__ Mt)
{
    __shared__ uint16_t tile[64][66];
    const int v0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int jj = ty; jj < 64; jj += 4) {
        const int j = j0 + jj, v = v0 + tx;
        tile[jj][tx] = (j < K && v < V) ? M[(size_t)j * V + v] : (uint16_t)0;
    }
    __syncthreads();
    for (int vv = ty; vv < 64; vv += 4) {
        const int v = v0 + vv, j = j0 + tx;
        if (v < V && j < K) Mt[(size_t)v * K + j] = tile[tx][vv];
    }
}

hipError_t launch_transpose_weights(const uint16_t *M, int K, int V, uint16_t *Mt, hipStream_t st)
{
    const dim3 grid((unsigned)((V + 63) / 64), (unsigned)((K + 63) / 64));
    transpose_weights_kernel<<<grid, 256, 0, st>>>(M, K, V, Mt);
    return hipGetLastError();
}

}  // namespace slimspec
