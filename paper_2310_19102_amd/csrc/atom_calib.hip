// Offline calibration for gfx950 (Section 5.1 of the paper): per-channel square sums of
// calibration activations and the reorder index that puts the channels with the highest
// square sums last.  A one-time cost; written for exactness and a unique result, not speed.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_internal.h"

namespace {

constexpr int kChunk = 256;               // rows per partial sum

// partial[chunk][k] = sum of x[t, k]^2 over the chunk's rows in ascending order (double).
// One thread per channel and chunk: consecutive threads read consecutive channels of a row.
__global__ __launch_bounds__(256)
void calib_partial_kernel(const __half *__restrict__ x, int64_t T, int64_t ldx, int K,
                          double *__restrict__ partial)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    const int64_t t0 = (int64_t)blockIdx.y * kChunk;
    const int64_t t1 = t0 + kChunk < T ? t0 + kChunk : T;
    double s = 0.0;
    for (int64_t t = t0; t < t1; ++t) {
        const double v = (double)__half2float(x[t * ldx + k]);
        s += v * v;
    }
    partial[(int64_t)blockIdx.y * K + k] = s;
}

// stat[k] = the chunk sums in ascending chunk order
__global__ __launch_bounds__(256)
void calib_total_kernel(const double *__restrict__ partial, int chunks, int K, double *__restrict__ stat)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += partial[(int64_t)c * K + k];
    stat[k] = s;
}

// idx[rank(i)] = i with rank(i) = number of channels before i in ascending (statistic,
// channel number) order: K comparisons per channel, every write goes to a different slot
__global__ __launch_bounds__(256)
void calib_rank_kernel(const double *__restrict__ stat, int K, int32_t *__restrict__ idx)
{
    __shared__ double tile[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const double si = i < K ? stat[i] : 0.0;
    int rank = 0;
    for (int j0 = 0; j0 < K; j0 += 256) {
        const int j = j0 + threadIdx.x;
        tile[threadIdx.x] = j < K ? stat[j] : 0.0;
        __syncthreads();
        const int n = K - j0 < 256 ? K - j0 : 256;
        for (int jj = 0; jj < n; ++jj) {
            const double sj = tile[jj];
            rank += (sj < si || (sj == si && j0 + jj < i)) ? 1 : 0;
        }
        __syncthreads();
    }
    if (i < K) idx[rank] = i;
}

}  // namespace

namespace atom_internal {

size_t calibrate_workspace_bytes(int64_t T, int K)
{
    const int64_t chunks = T > 0 ? (T + kChunk - 1) / kChunk : 0;
    return (size_t)(chunks + 1) * (size_t)K * sizeof(double);
}

hipError_t launch_calibrate_reorder(const void *x, int64_t T, int64_t ldx, int K, void *workspace,
                                    int32_t *idx, hipStream_t stream)
{
    const int chunks = (int)(T > 0 ? (T + kChunk - 1) / kChunk : 0);
    double *partial = static_cast<double *>(workspace);
    double *stat    = partial + (size_t)chunks * K;
    const unsigned kb = (unsigned)((K + 255) / 256);
    if (chunks > 0)
        hipLaunchKernelGGL(calib_partial_kernel, dim3(kb, (unsigned)chunks), dim3(256), 0, stream,
                           (const __half *)x, T, ldx, K, partial);
    hipLaunchKernelGGL(calib_total_kernel, dim3(kb), dim3(256), 0, stream, partial, chunks, K, stat);
    hipLaunchKernelGGL(calib_rank_kernel, dim3(kb), dim3(256), 0, stream, stat, K, idx);
    return hipGetLastError();
}

}  // namespace atom_internal
