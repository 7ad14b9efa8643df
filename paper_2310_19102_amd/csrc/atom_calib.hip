// Offline calibration for gfx950 (Section 5.1 of the paper): per-channel square sums of
// calibration activations and the reorder index that puts the channels with the highest
// square sums last.  A one-time cost; written for exactness (the sums are exact integers, whatever
// the order of the additions), not speed.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_internal.h"

namespace {

constexpr int kChunk = 256;               // rows per partial sum

// An exact square sum: the square of an fp16 value is an integer multiple of 2^-48 below 2^32, so a
// sum over up to 2^32 rows is an integer of at most 112 bits: two 64-bit words, any order.
struct U128 { unsigned long long lo, hi; };

__device__ __forceinline__ void add128(U128 &s, unsigned long long lo, unsigned long long hi)
{
    const unsigned long long t = s.lo + lo;
    s.hi += hi + (t < s.lo ? 1ull : 0ull);
    s.lo = t;
}

// x^2 in units of 2^-48 (Inf and NaN count as magnitude 2^16)
__device__ __forceinline__ void square_units(uint16_t h, unsigned long long &lo, unsigned long long &hi)
{
    const unsigned e = (h >> 10) & 31u, f = h & 1023u;
    const unsigned long long m = e == 0 ? f : (e == 31 ? 1024u : 1024u + f);     // |x| = m * 2^E
    const int E = e == 0 ? -24 : (e == 31 ? 6 : (int)e - 25);
    const unsigned long long m2 = m * m;                                         // < 2^22
    const int sh = 2 * E + 48;                                                   // 0 .. 60
    lo = m2 << sh;
    hi = sh > 0 ? m2 >> (64 - sh) : 0ull;
}

// partial[chunk][k] = exact sum of x[t, k]^2 over the chunk's rows.
// One thread per channel and chunk: consecutive threads read consecutive channels of a row.
__global__ __launch_bounds__(256)
void calib_partial_kernel(const uint16_t *__restrict__ x, int64_t T, int64_t ldx, int K,
                          U128 *__restrict__ partial)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    const int64_t t0 = (int64_t)blockIdx.y * kChunk;
    const int64_t t1 = t0 + kChunk < T ? t0 + kChunk : T;
    U128 s = {0ull, 0ull};
    for (int64_t t = t0; t < t1; ++t) {
        unsigned long long lo, hi;
        square_units(x[t * ldx + k], lo, hi);
        add128(s, lo, hi);
    }
    partial[(int64_t)blockIdx.y * K + k] = s;
}

// total[k] = sum of the chunk sums; stat[k] = the nearest double (ties to even) of total * 2^-48
__global__ __launch_bounds__(256)
void calib_total_kernel(const U128 *__restrict__ partial, int chunks, int K, U128 *__restrict__ total,
                        double *__restrict__ stat)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    U128 s = {0ull, 0ull};
    for (int c = 0; c < chunks; ++c) {
        const U128 p = partial[(int64_t)c * K + k];
        add128(s, p.lo, p.hi);
    }
    total[k] = s;
    double d;
    if (s.hi == 0) {
        d = (double)s.lo;                                   // (correctly rounded conversion)
    } else {
        // the top 64 bits with everything below folded into the lowest one, far below the
        // rounding position of the 64 -> 53 bit conversion
        const int sh = 64 - __clzll((long long)s.hi);       // 1 .. 48
        unsigned long long top = (s.hi << (64 - sh)) | (s.lo >> sh);
        if (s.lo & ((1ull << sh) - 1ull)) top |= 1ull;
        d = ldexp((double)top, sh);
    }
    stat[k] = ldexp(d, -48);
}

// idx[rank(i)] = i with rank(i) = number of channels before i in ascending (exact statistic,
// channel number) order: K comparisons per channel, every write goes to a different slot
__global__ __launch_bounds__(256)
void calib_rank_kernel(const U128 *__restrict__ total, int K, int32_t *__restrict__ idx)
{
    __shared__ U128 tile[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    U128 si = {0ull, 0ull};
    if (i < K) si = total[i];
    int rank = 0;
    for (int j0 = 0; j0 < K; j0 += 256) {
        const int j = j0 + threadIdx.x;
        U128 tj = {0ull, 0ull};
        if (j < K) tj = total[j];
        tile[threadIdx.x] = tj;
        __syncthreads();
        const int n = K - j0 < 256 ? K - j0 : 256;
        for (int jj = 0; jj < n; ++jj) {
            const U128 sj = tile[jj];
            const bool less  = sj.hi < si.hi || (sj.hi == si.hi && sj.lo < si.lo);
            const bool equal = sj.hi == si.hi && sj.lo == si.lo;
            rank += (less || (equal && j0 + jj < i)) ? 1 : 0;
        }
        __syncthreads();
    }
    if (i < K) idx[rank] = i;
}

}  // namespace

namespace atom_internal {

// [chunks][K] partial sums, [K] totals (16 bytes each), then [K] doubles
size_t calibrate_workspace_bytes(int64_t T, int K)
{
    const int64_t chunks = T > 0 ? (T + kChunk - 1) / kChunk : 0;
    return (size_t)(chunks + 1) * (size_t)K * sizeof(U128) + (size_t)K * sizeof(double);
}

hipError_t launch_calibrate_reorder(const void *x, int64_t T, int64_t ldx, int K, void *workspace,
                                    int32_t *idx, hipStream_t stream)
{
    const int chunks = (int)(T > 0 ? (T + kChunk - 1) / kChunk : 0);
    U128   *partial = static_cast<U128 *>(workspace);
    U128   *total   = partial + (size_t)chunks * K;
    double *stat    = reinterpret_cast<double *>(total + K);
    const unsigned kb = (unsigned)((K + 255) / 256);
    if (chunks > 0)
        hipLaunchKernelGGL(calib_partial_kernel, dim3(kb, (unsigned)chunks), dim3(256), 0, stream,
                           (const uint16_t *)x, T, ldx, K, partial);
    hipLaunchKernelGGL(calib_total_kernel, dim3(kb), dim3(256), 0, stream, partial, chunks, K, total, stat);
    hipLaunchKernelGGL(calib_rank_kernel, dim3(kb), dim3(256), 0, stream, total, K, idx);
    return hipGetLastError();
}

}  // namespace atom_internal
