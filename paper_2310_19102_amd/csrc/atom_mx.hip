// GEMM of the MX variant for gfx950: both operands hold FP4 E2M1 codes (normal channels) and
// FP8 E4M3 codes (outlier channels, last) with one E8M0 scale byte per block of 32 channels.
// The paper (Section 5.2, FP4 paragraph) expects hardware group scaling to take the
// dequantisation out of the kernel; on gfx950 that is v_mfma_scale_f32_32x32x64_f8f6f4, which
// multiplies each lane's 32 elements by 2^(scale byte - 127) inside the matrix core.  The
// K loop below is therefore nothing but operand movement and MFMAs.
//
// Operand layout of the instruction (checked on the hardware against a CPU sum):
//   A 32 x 64: lane l holds row l % 32; FP4: its 16 bytes are elements 32g .. 32g+31 of the
//     K = 64 step, g = l / 32, even element in the low nibble; FP8: its 32 bytes are elements
//     16g .. 16g+15 and 32+16g .. 32+16g+15.  B likewise with columns for rows.
//   scale: byte `op_sel` of the scale register of lane (row, g) is the scale of elements
//     32g .. 32g+31 of the row: for FP4 the lane's own 16 bytes, for FP8 the low (g = 0) or
//     high (g = 1) 16 bytes of both lanes of the row.  Either way an MX block of 32
//     consecutive channels has one scale.
//   C 32 x 32: lane l holds column l % 32, rows 8 (v / 4) + 4 (l / 32) + v % 4, v = 0..15.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "atom_gemm_common.h"
#include "atom_internal.h"

namespace {

typedef int   v4i  __attribute__((ext_vector_type(4)));
typedef int   v8i  __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256;         // workgroup tile
constexpr int NT = 512;                   // 8 wavefronts: 4 (rows of 64) x 2 (columns of 128)
constexpr int ROWB = 64;                  // bytes per tile row and K step: 128 FP4 or 64 FP8 channels
constexpr int STAGE = (BM + BN) * ROWB;   // 32 KB

struct MxParams {
    const uint8_t *a_q4, *a_q8, *a_e8;
    const uint8_t *w_q4, *w_q8, *w_e8;
    uint16_t *y;
    int64_t M, N, ldy;
    int K, O;
};

// 16-byte chunk `chunk` (0..3) of tile row `row`: rows r, r+4, r+8, r+12 would share a bank
// group (4 rows of 64 bytes span the 64 banks once), so the chunk index is rotated by row / 4;
// a fragment read (16 consecutive rows, one chunk index) and the loader's writes (4 rows x 4
// chunks per 16 lanes) then touch 16 different bank groups.
__device__ __forceinline__ int mx_lds_off(int row, int chunk)
{
    return row * ROWB + (((chunk + (row >> 2)) & 3) << 4);
}

template <int FMT, int OPSEL>
__device__ __forceinline__ v16f mfma_mx(v8i a, v8i b, v16f c, int sa, int sb)
{
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, FMT, FMT, OPSEL, sa, OPSEL, sb);
}

__device__ __forceinline__ v8i widen(v4i lo)
{
    return __builtin_shufflevector(lo, lo, 0, 1, 2, 3, -1, -1, -1, -1);
}
__device__ __forceinline__ v8i join(v4i lo, v4i hi)
{
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One K step per iteration: 64 bytes of every tile row, i.e. 128 FP4 channels (two MFMA
// sub-steps) or 64 FP8 channels (one).  Global -> registers -> LDS with two LDS stages:
// while step u is multiplied, step u+1 sits in the other stage and step u+2 is on its way
// into registers; one barrier per step.
__global__ __launch_bounds__(NT)
void mx_gemm_kernel(MxParams p)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, g = lane >> 5;

    const int tiles_m = (int)((p.M + BM - 1) / BM);
    const int bid = atom_gemm::xcd_contiguous_block_id();
    const int64_t m0 = (int64_t)(bid % tiles_m) * BM, n0 = (int64_t)(bid / tiles_m) * BN;

    const int K4 = p.K - p.O, NB = p.K >> 5;
    const int S4 = K4 >> 7, S8 = p.O >> 6, S = S4 + S8;

    // ---- loader: chunk id = tid + NT * i, row = id / 4 (A rows first), chunk = id % 4 = tid % 4;
    // 32-bit row numbers and offsets keep the addressing in few registers
    const int ch = tid & 3;
    uint32_t lrow[4];
    int dst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = (tid + NT * i) >> 2;                       // i < 2: A rows, else B rows
        int64_t r = i < 2 ? m0 + row : n0 + (row - BM);
        const int64_t last = (i < 2 ? p.M : p.N) - 1;
        lrow[i] = (uint32_t)(r < last ? r : last);                 // ragged tiles repeat the last row
        dst[i]  = mx_lds_off(row, ch);
    }
    auto fetch = [&](int u, uint4 (&v)[4]) {
        const bool f4 = u < S4;
        const uint32_t pitch = f4 ? (uint32_t)(K4 >> 1) : (uint32_t)p.O;
        const uint32_t col   = (uint32_t)(f4 ? u : u - S4) * ROWB + 16u * ch;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint8_t *base = i < 2 ? (f4 ? p.a_q4 : p.a_q8) : (f4 ? p.w_q4 : p.w_q8);
            v[i] = *reinterpret_cast<const uint4 *>(base + ((uint64_t)lrow[i] * pitch + col));
        }
    };
    auto stage = [&](int buf, const uint4 (&v)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(smem + buf * STAGE + dst[i]) = v[i];
    };

    // ---- scales: one dword (four blocks) per row and per FP4 step or pair of FP8 steps,
    // shifted at load time so that the lane's own block of a sub-step sits in byte 0 or 2
    uint32_t ea[2], eb[4];                                          // byte offsets of the rows' scale lines
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        int64_t r = m0 + 64 * wm + 32 * s + lr;
        r = r < p.M - 1 ? r : p.M - 1;
        ea[s] = (uint32_t)r * (uint32_t)NB;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        int64_t r = n0 + 128 * wn + 32 * t + lr;
        r = r < p.N - 1 ? r : p.N - 1;
        eb[t] = (uint32_t)r * (uint32_t)NB;
    }
    auto fetch_scales = [&](int u, int (&sa)[2], int (&sb)[4]) {
        // dword index of step u: FP4 step u -> u; FP8 steps 2j, 2j+1 -> S4 + j
        const uint32_t dw = 4u * (uint32_t)(u < S4 ? u : S4 + ((u - S4) >> 1));
#pragma unroll
        for (int s = 0; s < 2; ++s)
            sa[s] = (int)(*reinterpret_cast<const uint32_t *>(p.a_e8 + (ea[s] + dw)) >> (8 * g));
#pragma unroll
        for (int t = 0; t < 4; ++t)
            sb[t] = (int)(*reinterpret_cast<const uint32_t *>(p.w_e8 + (eb[t] + dw)) >> (8 * g));
    };

    v16f acc[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][t][v] = 0.0f;

    // fragment addresses: A rows 64 wm + 32 s + lr, B rows BM + 128 wn + 32 t + lr.  Rows 32
    // apart rotate alike, so sub-tiles are a constant 2048 bytes apart; chunk c + 2 is the
    // xor of chunk c's offset with 32.
    const int a_base = mx_lds_off(64 * wm + lr, g);
    const int b_base = mx_lds_off(BM + 128 * wn + lr, g);

    uint4 regs[4];
    int sa[2], sb[4], sa_nxt[2] = {0, 0}, sb_nxt[4] = {0, 0, 0, 0};
    fetch(0, regs);
    fetch_scales(0, sa, sb);
    stage(0, regs);
    if (S > 1) fetch(1, regs);
    __syncthreads();

    for (int u = 0; u < S; ++u) {
        const uint8_t *buf = smem + (u & 1) * STAGE;
        if (u + 1 < S) {
            stage((u + 1) & 1, regs);                     // that stage was last read in step u-1
            fetch_scales(u + 1, sa_nxt, sb_nxt);
        }
        if (u + 2 < S) fetch(u + 2, regs);

        if (u < S4) {
            // two sub-steps of 64 FP4 channels: bytes [0,32) and [32,64) of the row, the lane
            // takes chunk 2 k + g
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                v8i af[2], bf[4];
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    af[s] = widen(*reinterpret_cast<const v4i *>(buf + ((a_base ^ (32 * k)) + 2048 * s)));
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    bf[t] = widen(*reinterpret_cast<const v4i *>(buf + ((b_base ^ (32 * k)) + 2048 * t)));
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[s][t] = k == 0 ? mfma_mx<4, 0>(af[s], bf[t], acc[s][t], sa[s], sb[t])
                                           : mfma_mx<4, 2>(af[s], bf[t], acc[s][t], sa[s], sb[t]);
            }
        } else {
            // one step of 64 FP8 channels: the lane's low 16 bytes are chunk g (block 0 of the
            // step), its high 16 bytes chunk 2 + g (block 1); it carries the scale of block g,
            // byte 2 (u8 & 1) + g of the pair's dword.  Two halves of the columns at a time to
            // keep the fragments in few registers.
            const bool odd = (u - S4) & 1;
            v8i af[2];
#pragma unroll
            for (int s = 0; s < 2; ++s)
                af[s] = join(*reinterpret_cast<const v4i *>(buf + (a_base + 2048 * s)),
                             *reinterpret_cast<const v4i *>(buf + ((a_base ^ 32) + 2048 * s)));
#pragma unroll
            for (int th = 0; th < 2; ++th) {
                v8i bf[2];
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    bf[t] = join(*reinterpret_cast<const v4i *>(buf + (b_base + 2048 * (2 * th + t))),
                                 *reinterpret_cast<const v4i *>(buf + ((b_base ^ 32) + 2048 * (2 * th + t))));
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int t = 0; t < 2; ++t)
                        acc[s][2 * th + t] =
                            odd ? mfma_mx<0, 2>(af[s], bf[t], acc[s][2 * th + t], sa[s], sb[2 * th + t])
                                : mfma_mx<0, 0>(af[s], bf[t], acc[s][2 * th + t], sa[s], sb[2 * th + t]);
            }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) sa[s] = sa_nxt[s];
#pragma unroll
        for (int t = 0; t < 4; ++t) sb[t] = sb_nxt[t];
        __syncthreads();
    }

    // ---- store: lane holds column lr of sub-tile t, rows 8 (v / 4) + 4 g + v % 4 of sub-tile s
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t col = n0 + 128 * wn + 32 * t + lr;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + 64 * wm + 32 * s + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row < p.M && col < p.N)
                    p.y[row * p.ldy + col] = __half_as_ushort(__float2half_rn(acc[s][t][v]));
            }
        }
}

}  // namespace

namespace atom_internal {

hipError_t launch_mx_gemm(const void *a_q4, const void *a_q8, const void *a_e8, int64_t M,
                          const void *w_q4, const void *w_q8, const void *w_e8, int64_t N, int K,
                          int O, void *y, int64_t ldy, hipStream_t stream)
{
    MxParams p;
    p.a_q4 = (const uint8_t *)a_q4; p.a_q8 = (const uint8_t *)a_q8; p.a_e8 = (const uint8_t *)a_e8;
    p.w_q4 = (const uint8_t *)w_q4; p.w_q8 = (const uint8_t *)w_q8; p.w_e8 = (const uint8_t *)w_e8;
    p.y = (uint16_t *)y; p.M = M; p.N = N; p.ldy = ldy; p.K = K; p.O = O;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&mx_gemm_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE);
        if (err != hipSuccess) return err;
        attr_set = true;
    }
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    hipLaunchKernelGGL(mx_gemm_kernel, dim3((unsigned)tiles), dim3(NT), 2 * STAGE, stream, p);
    return hipGetLastError();
}

}  // namespace atom_internal
