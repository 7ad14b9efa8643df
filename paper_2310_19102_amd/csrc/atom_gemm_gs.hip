// Group GEMM for group sizes other than 128 (64 and 256: the group-size variation of Section
// 5.4.1 of the paper; arithmetic of Section 4.2, steps 1-3).
//
// Written for exactness and plainness, not speed (the tuned kernels are built around the group
// of 128 of the paper's set-up, Section 5.1): a workgroup of four wavefronts owns a 64 x 64 tile,
// a wavefront a 32 x 32 tile of the INT8 MFMA 32x32x32.  Fragments come straight from global
// memory (a lane holds one operand row's 16 bytes of the current K chunk), INT4 codes widened to
// the high halves of bytes (16 * code, both operands: the integer sum is 256 * P, the 2^-8 folded
// into the weight scale).  Per group g, in ascending order as the oracle does it:
//   P = sum over the group's channels (int32, exact);  acc = fmaf(float(P), as[m,g] * ws[n,g], acc)
// so Y is the oracle's Y bit for bit.
//
// MFMA 32x32x32 i8: lane l supplies row (l & 31) of its operand and the 16 bytes of K chunk
// (l >> 5); the result has column (l & 31) in lane l and rows 8*(r>>2) + 4*(l>>5) + (r&3) in
// register r = 0..15.  Activations are the row operand.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_gemm_common.h"
#include "atom_internal.h"

namespace {

using namespace atom_gemm;

typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4i nib_lo(uint4 w)
{
    v4u t = {(w.x << 4) & 0xF0F0F0F0u, (w.y << 4) & 0xF0F0F0F0u, (w.z << 4) & 0xF0F0F0F0u, (w.w << 4) & 0xF0F0F0F0u};
    return __builtin_bit_cast(v4i, t);
}
__device__ __forceinline__ v4i nib_hi(uint4 w)
{
    v4u t = {w.x & 0xF0F0F0F0u, w.y & 0xF0F0F0F0u, w.z & 0xF0F0F0F0u, w.w & 0xF0F0F0F0u};
    return __builtin_bit_cast(v4i, t);
}

__global__ __launch_bounds__(256)
void w4a4_gemm_gs_kernel(const GemmParams p, int gs)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, c = lane >> 5;
    const int K4 = p.K - p.O, G = p.K / gs, G4 = K4 / gs;
    const int64_t m0 = (int64_t)blockIdx.y * 64 + (wave >> 1) * 32;
    const int64_t n0 = (int64_t)blockIdx.x * 64 + (wave & 1) * 32;
    // operand rows of this lane (clamped: rows past the end are computed and never stored)
    const int64_t ma = min(m0 + r, p.M - 1), nb = min(n0 + r, p.N - 1);
    const uint8_t *a4 = p.a_q4 + ma * (K4 >> 1) + c * 16, *w4 = p.w_q4 + nb * (K4 >> 1) + c * 16;
    const int8_t  *a8 = p.a_q8 + ma * p.O + c * 16, *w8 = p.w_q8 + nb * p.O + c * 16;
    const uint16_t *ws = p.w_scale + nb * G;         // the lane's output column
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

    for (int g = 0; g < G; ++g) {
        v16i P;
#pragma unroll
        for (int i = 0; i < 16; ++i) P[i] = 0;
        const bool is4 = g < G4;
        if (is4) {
            // 64 channels per trip: 32 bytes of a row, two K chunks of 16 bytes
            for (int t = 0; t < gs / 64; ++t) {
                const size_t off = ((size_t)g * gs + (size_t)t * 64) >> 1;
                const uint4 a = *reinterpret_cast<const uint4 *>(a4 + off);
                const uint4 w = *reinterpret_cast<const uint4 *>(w4 + off);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(nib_lo(a), nib_lo(w), P, 0, 0, 0);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(nib_hi(a), nib_hi(w), P, 0, 0, 0);
            }
        } else {
            for (int t = 0; t < gs / 32; ++t) {
                const size_t off = (size_t)(g - G4) * gs + (size_t)t * 32;
                const v4i a = *reinterpret_cast<const v4i *>(a8 + off);
                const v4i w = *reinterpret_cast<const v4i *>(w8 + off);
                P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, w, P, 0, 0, 0);
            }
        }
        const float wsf = half_bits_to_float(ws[g]) * (is4 ? (1.0f / 256.0f) : 1.0f);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t m = m0 + 8 * (i >> 2) + 4 * c + (i & 3);
            const int64_t mc = m < p.M ? m : p.M - 1;
            const float sa = half_bits_to_float(p.a_scale[mc * G + g]);
            acc[i] = fmaf((float)P[i], sa * wsf, acc[i]);
            if (p.partials && m < p.M && n0 + r < p.N)
                p.partials[(m * p.N + (n0 + r)) * G + g] = is4 ? P[i] >> 8 : P[i];     // 256 * P: exact shift
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t m = m0 + 8 * (i >> 2) + 4 * c + (i & 3);
        if (m < p.M && n0 + r < p.N) p.y[m * p.ldy + n0 + r] = __half_as_ushort(__float2half_rn(acc[i]));
    }
}

}  // namespace

namespace atom_internal {

hipError_t launch_w4a4_gemm_gs(const GemmArgs &a, int group_size, hipStream_t stream)
{
    GemmParams p;
    p.a_q4 = a.a_q4; p.a_q8 = a.a_q8; p.a_scale = a.a_scale;
    p.w_q4 = a.w_q4; p.w_q8 = a.w_q8; p.w_scale = a.w_scale;
    p.y = a.y; p.partials = a.partials;
    p.M = a.M; p.N = a.N; p.ldy = a.ldy; p.K = a.K; p.O = a.O;
    const dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64));
    hipLaunchKernelGGL(w4a4_gemm_gs_kernel, grid, dim3(256), 0, stream, p, group_size);
    return hipGetLastError();
}

}  // namespace atom_internal
