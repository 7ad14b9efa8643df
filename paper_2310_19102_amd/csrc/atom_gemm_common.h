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

// Byte offset of 16-byte chunk `chunk` (0..7) of tile row `row` (128 bytes per row).
// Measured on gfx950: a 128-bit LDS read is served 16 lanes per pass out of 64 banks of
// 4 bytes, so two consecutive rows span the banks once, and a fragment read (16
// consecutive rows, one chunk index) is conflict-free only if those rows land on 16
// different 16-byte bank groups.  Xor-ing the chunk with the low three row bits alone
// repeats after eight rows (2-way conflicts, half the read rate); folding row bit 3 in
// separates rows r and r+8.  The loader's 128-bit writes (4 rows x 4 chunks per 16
// lanes) run at their full rate with it as well.  The pattern has period 16 rows.
__device__ __forceinline__ int lds_off(int row, int chunk)
{
    return row * 128 + (((chunk ^ row ^ ((row >> 3) & 1)) & 7) << 4);
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
// The same on weight codes re-tiled by launch_tile_weight (w_q4, w_q8 of p are the tiled arrays).
hipError_t launch_tile_weight(const void *q4, const void *q8, int64_t N, int K, int O, void *t4, void *t8,
                              hipStream_t stream);
bool decode_tiled_supported(const GemmParams &p);
// rounds of workgroups (one per CU) the streaming kernels take for more than 64 rows
int decode_rounds(const GemmParams &p);
hipError_t launch_decode_tiled(const GemmParams &p, hipStream_t stream);

}  // namespace atom_gemm
#endif
