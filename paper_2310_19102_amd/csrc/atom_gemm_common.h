// Shared definitions of the group-GEMM kernels.
#ifndef ATOM_GEMM_COMMON_H
#define ATOM_GEMM_COMMON_H

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace atom_gemm {

typedef int v4i  __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmParams {
    const uint8_t *a_q4; const int8_t *a_q8; const uint16_t *a_scale;
    const uint8_t *w_q4; const int8_t *w_q8; const uint16_t *w_scale;
    uint16_t *y; int32_t *partials;
    int64_t M, N, ldy;
    int K, O;
};

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return __half2float(__ushort_as_half(h));
}

// Byte offset of 16-byte chunk `chunk` (0..7) of tile row `row`; the xor keeps
// eight consecutive rows on eight different bank groups.
__device__ __forceinline__ int lds_off(int row, int chunk)
{
    return row * 128 + (((chunk ^ row) & 7) << 4);
}


// Logical tile index of this workgroup.  Hardware deals consecutive workgroup
// ids round-robin to the 8 XCDs; give every XCD a contiguous run of logical
// tiles so neighbouring tiles (which share operand rows) meet in one L2.
__device__ __forceinline__ int xcd_contiguous_block_id()
{
    const int nb = gridDim.x, b = blockIdx.x;
    const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
    return xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
}

// Big-tile kernel for compute-bound sizes, M > 64 (atom_gemm_big.hip).
hipError_t launch_big(const GemmParams &p, hipStream_t stream);

// Weight-streaming kernel for decode-sized M <= 64 (atom_gemm_decode.hip).
hipError_t launch_decode(const GemmParams &p, hipStream_t stream);

}  // namespace atom_gemm
#endif
